"""MI355X-native cached denoising step of a DeepCache-style video UNet (LightCache hot path).

`binding` forwards to liblightcache.so (hand-written HIP for gfx950); `synth` draws the seeded
synthetic inputs; `build` compiles the library.
"""
