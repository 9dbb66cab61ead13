"""MI355X-native gradient compressor (accumulate -> Top_k / Gaussian_k select -> compact ->
residual).  `sparsify` is the binding over the HIP library; `synth` makes seeded inputs."""
