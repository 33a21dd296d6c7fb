"""MI355X-native product-quantization ADC scan (hand-written HIP behind a C ABI).

``datagen`` holds the seeded input generators; ``binding`` is the thin Python
layer over ``libpqadc.so`` (argument marshalling only).
"""
__all__ = ["datagen", "binding"]
