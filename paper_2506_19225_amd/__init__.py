"""MI355X-native chunk-based pre-filling attention and bi-level KV decoding (Video-XL-2,
"Efficiency Optimization").  `vxl` is the ctypes binding of the C-ABI HIP library;
`workloads` holds the seeded synthetic inputs.  Nothing is loaded at package import."""
