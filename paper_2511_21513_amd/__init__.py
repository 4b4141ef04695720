"""MI355X-native fused integer attention (IntAttention hot path).

``paper_2511_21513_amd.binding`` wraps the C-ABI library (``include/intattn.h``).  Importing the
package loads nothing native; the binding loads the HIP library on first use and
raises if it has not been built.
"""
__all__ = ["binding", "build"]
