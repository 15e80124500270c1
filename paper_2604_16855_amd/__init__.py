"""MI355X-native DSTG + DCRP W4A4 quantized linear (COD-TDQ hot path).

`paper_2604_16855_amd.tdq` is the thin binding over the C-ABI library
(`libtdq.so`, hand-written HIP for gfx950); `paper_2604_16855_amd.inputs`
holds the seeded synthetic input generators.  Importing the package loads
neither torch nor the library; `tdq` does both on first use.
"""
__all__ = ["inputs", "tdq"]
