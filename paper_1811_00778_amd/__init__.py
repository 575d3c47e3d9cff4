"""MI355X-native hot path of HCNN's encrypted CNN inference (RNS-form FV arithmetic).

Import `paper_1811_00778_amd.binding` for the GPU entry points; nothing here falls
back to a CPU implementation.
"""
__all__ = ["binding", "layers", "build"]
