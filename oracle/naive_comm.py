"""The back-of-envelope communication volumes of the worked example in Sec. 2.2
(five 300-wide FC layers, batch 400, 16 GPUs, 4-byte elements).  This is the
paper's *simple* formula (size x devices x 2), not the k-cut cost model."""


def param_bytes(width, layers, elem=4):
    return width * width * layers * elem


def activation_bytes(batch, width, layers, elem=4):
    return batch * width * layers * elem


def data_parallel(width, layers, n_dev, elem=4):
    # gather every device's gradients, then send the updated parameters back
    return param_bytes(width, layers, elem) * n_dev * 2


def model_parallel(batch, width, layers, n_dev, elem=4):
    # activations forward and their gradients backward
    return activation_bytes(batch, width, layers, elem) * n_dev * 2


def hybrid_across(width, layers, groups, elem=4):
    # data parallelism across the groups: every group's gradients gathered, the parameters sent back
    return param_bytes(width, layers, elem) * groups * 2


def hybrid_within(batch, width, layers, groups, per_group, elem=4):
    # model parallelism inside one group, on that group's share of the batch
    return activation_bytes(batch, width, layers, elem) // groups * per_group * 2


def hybrid(batch, width, layers, groups, per_group, elem=4):
    return hybrid_across(width, layers, groups, elem) + groups * hybrid_within(batch, width, layers, groups, per_group, elem)
