"""The scheduler's test instances (workloads/lda.py) as the scheduler's own Model / Device objects."""
from workloads.lda import FORMATS, hand_model, random_instance  # noqa: F401  (re-exported for the tests)


def as_objects(model, devices):
    from paper_2504_08791_amd import halda
    mo = halda.Model(L=model["L"], flops=dict(model["flops"]), flops_out=dict(model["flops_out"]), b=model["b"], b_i=model["b_i"],
                     b_o=model["b_o"], V=model["V"], kv_bytes_per_token=model["kv"], n_kv=model["n_kv"], c_cpu=model["c_cpu"], c_gpu=model["c_gpu"])
    ds = [halda.Device(name=f"d{m}", os=d["os"], gpu=d["gpu"], uma=d["uma"], d_avail=d["d_avail"], d_gpu_avail=d["d_gpu_avail"],
                       d_swapout=d["swap_cap"], s_disk=d["s_disk"], s_cpu=dict(d["s_cpu"]), s_gpu=dict(d["s_gpu"]), T_cpu=d["T_cpu"],
                       T_gpu=d["T_gpu"], t_kv_cpy_cpu=d["t_kv_cpy_cpu"], t_kv_cpy_gpu=d["t_kv_cpy_gpu"], t_ram_vram=d["t_ram_vram"],
                       t_vram_ram=d["t_vram_ram"], t_comm=d["t_comm"]) for m, d in enumerate(devices)]
    return mo, ds
