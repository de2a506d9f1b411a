"""MI355X-native scoring path of MaaSO's placer and distributor (gfx950 HIP kernels + C-ABI)."""
