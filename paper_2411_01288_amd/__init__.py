"""MI355X-native expert-specific MoE FFN layer (HEXA-MoE operators), C-ABI + thin binding.

Importing the package does not load the HIP library; `paper_2411_01288_amd.binding`
does, and raises if it is missing.
"""
