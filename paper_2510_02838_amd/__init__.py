"""MI355X-native Diffuse stage (diffusion-transformer denoising loop): HIP kernels behind a
C ABI (include/dit.h), with a ctypes binding of the same names in `binding`."""
