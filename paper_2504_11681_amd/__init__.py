"""tfno: fused FNO spectral convolution (TurboFNO, arxiv 2504.11681) for AMD MI355X (gfx950).

The compute path is the HIP library ``libtfno.so`` (C ABI declared in
``include/tfno.h``); ``binding`` marshals PyTorch device pointers into it.
Nothing here falls back to the CPU: without the built library every call raises.
"""
__all__ = ["binding", "inputs"]
