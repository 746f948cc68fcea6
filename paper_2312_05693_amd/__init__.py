"""agq: the W4A8 / W4A4 quantized linear layer of Agile-Quant (arxiv 2312.05693)
as HIP kernels for MI355X behind a C ABI (include/agq.h).

`binding` wraps the C ABI (needs the built libagq.so and torch); `synth` draws
the seeded synthetic inputs; `build` compiles the library with hipcc."""
