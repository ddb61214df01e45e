"""MI355X-native hot path of TIDE: the per-denoise-step MoE expert layer against a
GPU-resident expert cache, the interval hit counter and the top-B refresh.

`binding` mirrors the C ABI of include/tide.h one to one; `build` compiles libtide.so."""
