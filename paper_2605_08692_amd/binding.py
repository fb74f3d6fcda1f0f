"""placeholder"""
class AaacError(RuntimeError): pass
NVFP4, INT4 = 0, 1
def _todo(*a, **k): raise AaacError("not built")
aaac_act_stats = aaac_act_stats_workspace = aaac_dequant = aaac_encode = aaac_fit = aaac_fit_batch = aaac_fit_workspace = library = library_path = _todo
