from workloads.harness import DeviceLayer, HostLayer, err_metric, to_device  # noqa: F401
