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


def hybrid(batch, width, layers, groups, per_group, elem=4):
    across = param_bytes(width, layers, elem) * groups * 2
    within = activation_bytes(batch, width, layers, elem) // groups * per_group * 2
    return across + groups * within
