"""MI355X-native PrecisionBatching hot path (bit-decomposed quantized matrix product).

The HIP library is loaded lazily on the first call into `paper_2003_00822_amd.pb`;
importing the package (e.g. for `synth`) does not need it.
"""
